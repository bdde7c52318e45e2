"""MI355X-native block-level attention for one FCP worker (C-ABI library + thin binding)."""
