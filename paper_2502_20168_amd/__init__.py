"""MI355X-native resettable S5 scan layer (forward + gradient pass) behind a C-ABI library.

`workloads` draws the synthetic inputs; `binding` marshals torch tensors into the C-ABI calls of
libssmscan.so.  The HIP library is loaded lazily on first use and its absence is an error: there
is no CPU fallback.
"""
