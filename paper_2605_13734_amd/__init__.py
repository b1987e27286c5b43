"""MI355X-native KV-cache compress / decompress path (KVServe, section 5.1: Q and C stages).

`kvc`  : thin ctypes binding of the C-ABI library (HIP kernels for gfx950)
`kvgen`: seeded synthetic KV generator
Importing this package loads nothing; `kvc.load()` fails loudly if the library is not built.
"""
