"""CPU oracle for the CacheCard hot path.  Test infrastructure only: see qkv_ref.cpp."""
