"""MI355X-native implementation of one device's share of an Astra attention layer.

``workloads`` (seeded synthetic inputs) needs numpy only.  The compute entry
points live in ``binding`` and call the HIP library through its C ABI; they
raise if the library has not been built -- there is no CPU fallback.
"""
