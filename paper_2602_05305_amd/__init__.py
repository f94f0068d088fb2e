"""FlashBlock attention hot path for MI355X (gfx950): Python binding over libflashblock.so."""
