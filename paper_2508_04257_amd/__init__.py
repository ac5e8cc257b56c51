"""MI355X-native hot path of KVSink: sink prediction, sink-preserving low-bit KV-cache
quantisation and decode attention over the packed cache (hand-written HIP for gfx950 behind
a small C ABI).  ``binding`` loads the shared library on first use and raises if it is not
built; nothing here computes on the CPU."""
