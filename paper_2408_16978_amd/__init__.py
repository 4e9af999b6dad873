"""MI355X-native chunked causal attention (forward + backward, with host
offload of key/value chunks): thin Python binding over the C-ABI HIP library."""
