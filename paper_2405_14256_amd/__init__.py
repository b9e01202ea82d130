"""MI355X-native hot path of ZipCache (arXiv 2405.14256): probe saliency,
salient-token selection, mixed-precision quantize-and-pack, and single-query
attention over the packed cache.  All arithmetic runs in the HIP library
(`libzipcache.so`); this package only marshals arguments."""

__all__ = ["binding", "probes", "workloads"]
