"""MI355X-native hot path of Memo (arXiv 2407.12117): causal attention fwd/bwd and
token-wise activation swap behind the C-ABI library libmemo.so."""
