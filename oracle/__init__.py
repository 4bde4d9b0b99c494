"""TEST INFRASTRUCTURE ONLY -- the slow CPU oracle (see nature_cnn.py)."""
