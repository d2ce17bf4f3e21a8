"""libgbmuf: the random-gossip BMUF synchronisation step (arXiv 1909.09010, Algorithm 1) for
AMD MI355X.  ``binding`` wraps the C ABI of ``include/gbmuf.h``; ``workloads`` holds the
seeded synthetic parameter sets (shapes and value distributions only, no arithmetic of the
method).  Importing ``binding`` fails if ``libgbmuf.so`` has not been built."""
