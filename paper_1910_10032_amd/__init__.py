"""MI355X-native batched WFST Viterbi decoder: Python binding of the C-ABI library."""
