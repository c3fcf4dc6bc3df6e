"""MI355X-native embedding-cache step (lookup / update / flush with per-embedding clocks).

`hetcache` is the thin ctypes binding over the C-ABI library built from `csrc/`;
`workloads` holds the seeded synthetic input generators.  The library is loaded lazily, so
importing this package needs neither a GPU nor a built extension.
"""
__all__ = ["workloads", "hetcache"]
