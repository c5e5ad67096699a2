"""Head-wise MMDiT joint attention (full / arrow / output-cache per head) for MI355X."""
