"""CPU oracle for the FreeKV retrieval-decode path (test infrastructure only)."""
