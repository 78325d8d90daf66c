"""CPU oracle (test infrastructure only; the GPU package never imports this)."""
