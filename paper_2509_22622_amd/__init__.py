"""MI355X-native sink+window attention over a rolling KV cache (LongLive hot path).

The compute lives in the HIP library behind the C-ABI declared in
``include/longlive.h``; :mod:`.binding` marshals arguments to it and nothing else.
Importing this package does not load the library; :func:`binding.lib` does.
"""
