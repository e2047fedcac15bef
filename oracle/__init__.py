"""CPU oracle (test infrastructure only; see rectify_router.py)."""
